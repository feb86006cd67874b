"""CPU ORACLE -- test infrastructure, not the product.

A plain, slow, obviously-correct CPU evaluation of what one Sync EASGD round
computes (paper Eq. (1), (2), (5), (6); Section 5.1 steps (1)-(5)).  It is the
yardstick the HIP library is compared against and shares no code with it.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.

* ``oracle.elastic``  -- exchange-and-update (C, double arithmetic, fp32 storage); also the
  synchronous data-parallel SGD round on replicas (Section 2.3, Section 6.2; Eq. (3),(4)) and the master
  serving one worker at a time (Algorithm 1; Async EASGD / Async MEASGD of Section 5.1)
* ``oracle.elastic_bf16`` -- the same update with gradients and momentum buffers stored as bfloat16
  (an extension; numpy; the stored 16-bit code is decided in fp32, the rest in double)
* ``oracle.mlp_grad`` -- per-worker minibatch gradient of a dense ReLU MLP with
  softmax cross-entropy (numpy, double arithmetic)
"""
from .elastic import (async_easgd, build, easgd_round, measgd_round, num_threads, set_num_threads,  # noqa: F401
                      sync_sgd_round)
from .elastic_bf16 import bf16_round, bf16_widen, easgd_round_bf16, measgd_round_bf16  # noqa: F401
from .mlp_grad import mlp_grad, mlp_grad_all_workers, layer_slices  # noqa: F401
