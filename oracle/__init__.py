"""CPU oracle for the LRQ-DiT quantized linear layer (numpy, fp64).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the
HIP path is checked against; it is imported by tests/, by the smoke check and by
the benchmark's cpu_baseline leg, never by the product path.  It shares no code,
table or constant with the HIP sources and does not import the GPU package.

What follows the paper and where:

* rotation.py  - Sylvester Hadamard matrix and its butterfly form
                 (Preliminaries, "Rotation Transformation", Eq. hadamard), the
                 dense rotation X.R used for the outlier-aware branch of the
                 Adaptive Rotation Scheme (Method, ARS case equation), that branch in
                 its structured form X.R1.P.R2 (block-diagonal rotations, staggered
                 permutation) and the greedy builder of R1, P, R2 from calibration
                 activations (equation R^i = E R~ Q E).
* calib.py     - fluctuation metric J and the threshold rule that picks a layer's
                 rotation (Method, Eq. J and the ARS case equation); per-channel
                 smoothing factor (Experiment, "Implementation Details").
* actquant.py  - per-token dynamic uniform quantizer (Preliminaries, Eq. 1, in
                 its symmetric absmax form; Experiment, "Implementation Details":
                 per-token dynamic activations).
* tlq.py       - Twin-Log Quantization: log2 transform, sign masks, twin
                 clamp-round quantizers (Eq. log-based quantizer), search-based
                 clipping (Eq. hyperparameters clip), dequantization (Eq. dequant),
                 exponent split and integerisation ("Hardware Implementation").
* fp8.py       - FP8 E4M3 conversion (the operand format of the FP8 value map: levels with I = 3 mantissa bits).
* qlinear.py   - the quantized linear layer Y = s_x * s_w * (I_x . I_w) assembled
                 from the above (last equation of "Hardware Implementation").

Pins (tests/test_oracle_*.py) and what is parity-unpinned by the paper: the int8
normalisation of the level table and the [1, 2^(b-1)] clamp of the negative twin
are this build's readings of points the paper leaves open; they are pinned only
by their own stated definitions, everything else against closed forms, library
special cases and brute force.  The greedy rotation builder fills in what the paper
leaves unnamed (which matrix initialises R~, which Q, how c* is chosen, the dealing
order of the staggered permutation); it is pinned by the printed matrix product, by
orthogonality and by the Lemma's ||x'||_inf = ||x||_inf / sqrt(C) on a single outlier,
and is otherwise parity-unpinned by the paper.  The smoothing factor's formula is the
cited SmoothQuant one (the paper only names the migration strength).
"""
from .bf16 import bf16_bits_to_f64, f64_to_bf16_bits  # noqa: F401
from .rotation import (hadamard_matrix, fwht_blocks, rotate_hadamard, rotate_dense, rotate_blockdiag,  # noqa: F401
                       rotate_blockperm, zigzag_permutation, greedy_block_rotation, build_outlier_rotation)
from .calib import fluctuation_J, select_rotation, smoothing_factor, smooth_weights  # noqa: F401
from .actquant import quantize_per_token, quantize_per_token_asym, pack_act_codes4, unpack_act_codes4  # noqa: F401
from .tlq import (TLQParams, tlq_calibrate, tlq_encode, tlq_exponents, tlq_dequant,  # noqa: F401
                  tlq_level_values, tlq_lut, tlq_lut_fp8, pack_codes, unpack_codes)
from .fp8 import e4m3_bits_to_f64, f64_to_e4m3_bits  # noqa: F401
from .qlinear import (ars_rotate_quant, ars_rotate_quant_asym, qlinear, qlinear_from_parts,  # noqa: F401
                      qlinear_from_parts_asym, qlinear_levels_from_parts, qlinear_fp8_from_parts, act_codes_to_e4m3,
                      reference_linear)
