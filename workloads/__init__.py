"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This package only *draws* inputs (graphs, query batches, negatives, initial
parameter values).  It contains none of the method's arithmetic: no operator,
score, loss, gradient, optimiser or planning code lives here, so that the
oracle and the HIP library stay independent of each other.
"""
from .configs import CONFIGS, Config, get_config, TEMPLATES, ALL14, EPFO9  # noqa: F401
from .kg import KG, make_kg  # noqa: F401
from .queries import QueryBatch, make_batch, make_negatives, batch_from_trees  # noqa: F401
from .params import (make_params, make_box_params, make_sem_features, PARAM_NAMES, MLP_PARAM_NAMES,  # noqa: F401
                     BOX_PARAM_NAMES)  # noqa: F401
