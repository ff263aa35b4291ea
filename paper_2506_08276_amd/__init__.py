"""MI355X-native hot path of LEANN's search (arXiv 2506.08276): ctypes binding of libleann.so."""
from .binding import *  # noqa: F401,F403
from .binding import (LeannError, load_library, leann_create, leann_destroy, leann_embed, leann_build_pq,  # noqa: F401
                      leann_pq_export, leann_pq_import, leann_pq_wrap, leann_pq_info, leann_pq_free, leann_adc,
                      leann_search, leann_search_updates, leann_build_graph, leann_top_degree, leann_set_limits, leann_profile_begin, leann_profile_end, EXPORTS, LIB_PATH)
