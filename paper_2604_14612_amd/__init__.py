"""MI355X-native self-speculative decoding hot path (ConfLayers): Python binding of libssd.so."""
from .binding import (Context, Search, SsdError, lib, make_config, pack_weights, search_defaults, select_defaults,
                      ssd_hbm_read_probe, ssd_select_skip, ssd_uniform_skip, SYMBOLS, LIB_PATH,
                      SSD_OK, SSD_EINVAL, SSD_ESTATE, SSD_ECAPACITY, SSD_ENOMEM, SSD_EHIP, SSD_MAX_K,
                      SSD_PREFILL_ROWS)
from .generate import generate_conflayers, generate_vanilla

__all__ = ["Context", "Search", "SsdError", "lib", "make_config", "pack_weights", "search_defaults", "select_defaults",
           "ssd_hbm_read_probe", "ssd_select_skip", "ssd_uniform_skip", "SYMBOLS", "LIB_PATH",
           "SSD_OK", "SSD_EINVAL", "SSD_ESTATE", "SSD_ECAPACITY", "SSD_ENOMEM", "SSD_EHIP", "SSD_MAX_K",
           "SSD_PREFILL_ROWS", "generate_conflayers", "generate_vanilla"]
