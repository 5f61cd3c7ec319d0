"""Profiling-metric study: the paper's metric-selection procedure (Sec. 2.3, Alg. 1-2) applied to
rocprofv3 hardware counters of this library's own kernel variants on MI355X.

    python -m paper_2511_01884_amd.metric_study.collect  OUT_DIR     # runs rocprofv3, writes CSV dumps
    python -m paper_2511_01884_amd.metric_study.analyse  OUT_DIR REPORT.md

Tasks are operator shapes; the kernels of a task are the tiled kernel's tile shapes and modes
(128/256 tiles, one or two workgroups per compute unit, fused or two-pass), all computing the same
result.  The paper draws 100 generated kernels per task and keeps the 5 fastest and 5 slowest
(Alg. 1); here every variant the library has is used.
"""
