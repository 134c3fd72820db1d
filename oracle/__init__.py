"""WKV6 prefill oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the GPU library
and never imports it.

``wkv6_oracle``   sequential fp64 recurrence in plain C (``wkv6_oracle.c``),
                  threaded over (batch, head) units.
``wkv6_numpy``    an independent NumPy fp64 twin of the same recurrence
                  (``wkv6_numpy.py``), used to cross-check the C build.
``finch_c2_oracle`` / ``finch_c2_numpy``
                  the Finch-C2 form of the time mix (key times one minus the decay, second
                  value added to the read-out, no bonus), ``finch_c2_oracle.c`` and its twin.
``key_compress_oracle``
                  the GOLD key compression c_t = x_t W^KD as three plain loops
                  (``key_compress_oracle.c``).
``layernorm_heads_numpy`` / ``head_moments_numpy``
                  the LayerNorm over the concatenated heads of the Finch-C2 output equation and
                  the per-head partial moments it can be combined from (``layernorm_numpy.py``).
``lora_numpy`` / ``decay_logits_numpy``
                  the low-rank operator lambda + tanh(x A) B and its last factor, the decay logits
                  from y = tanh(. A) (``decay_lora_numpy.py``).
``lerp_numpy`` / ``token_shift_numpy`` / ``ddlerp_numpy`` / ``decay_lora_input_numpy``
                  the operators in front of the decay path: token shift, ddlerp with its inner lora,
                  and y = tanh(ddlerp_d(x_t, x_{t-1}) A_omega) (``ddlerp_numpy.py``).
"""
from .cbuild import build_oracle, finch_c2_oracle, key_compress_oracle, wkv6_oracle  # noqa: F401
from .ddlerp_numpy import decay_lora_input_numpy, ddlerp_numpy, lerp_numpy, token_shift_numpy  # noqa: F401
from .decay_lora_numpy import decay_logits_numpy, lora_numpy  # noqa: F401
from .layernorm_numpy import head_moments_numpy, layernorm_heads_numpy  # noqa: F401
from .wkv6_numpy import finch_c2_numpy, wkv6_numpy  # noqa: F401
