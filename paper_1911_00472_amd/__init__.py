"""MI355X (gfx950) decoder for Progressive Compressed Records: C-ABI library in csrc/ built to
libpcr.so, plus a thin ctypes binding with the same entry-point names."""
from .binding import (E_ARG, E_DEVICE, E_FORMAT, E_NOMEM, E_RANGE, E_TRUNCATED, E_UNSUPPORTED, LIB_PATH, NUM_STAGES, OK,
                      STAGE_NAMES, SYMBOLS, Loader, PcrError, Record, lib, pcr_open, pcr_open_device, prefix_length,
                      probe_scalar_issue_rate, record_write, record_write_indexed, scan_ends, transcode_files, transcode_progressive, transcode_symbol_counts)

__all__ = ["Record", "Loader", "prefix_length", "scan_ends", "record_write", "record_write_indexed", "transcode_progressive", "transcode_symbol_counts", "transcode_files", "pcr_open", "pcr_open_device", "probe_scalar_issue_rate", "PcrError", "lib", "SYMBOLS", "LIB_PATH", "STAGE_NAMES", "NUM_STAGES",
           "OK", "E_ARG", "E_FORMAT", "E_TRUNCATED", "E_UNSUPPORTED", "E_RANGE", "E_NOMEM", "E_DEVICE"]
