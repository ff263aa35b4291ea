"""Seeded synthetic inputs shared by the oracle-side and GPU-side harnesses.

Holds none of the method's arithmetic (no encoder, no PQ, no search): only
random weights, token stores, and graph fixtures built from a given embedding
matrix.  Everything is a deterministic function of its seed.
"""
from .configs import TINY, BASE, SMALL, BASE_S128, SEED0, config_seed  # noqa: F401
from .weights import encoder_weights, weight_layout, to_bf16_exact  # noqa: F401
from .chunks import (uniform_chunks, topic_chunks, make_topics, family_corpus, family_queries,  # noqa: F401
                     make_latent_space, latent_corpus, latent_queries)  # noqa: F401
from .graphs import knn_graph, navigable_fixture, to_csr, add_ring, max_in_degree_node, hub_slots  # noqa: F401
