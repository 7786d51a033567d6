"""CPU oracle of the compressed CDC shuffle (test infrastructure only).

Nothing in the GPU product path may import this package; it exists so that
tests, the smoke check and the benchmark's CPU-baseline leg have an
independent answer to compare with.
"""
from .ccdc_oracle import (  # noqa: F401
    CompressionPlan,
    OraclePlan,
    build_library,
    build_plan,
    closed_form_elems,
    combine,
    combine_h32,
    decode,
    decode_h32,
    direct,
    direct_h16,
    encode,
    encode_h32,
    h16_narrow,
    h16_widen,
    label_rank,
    map_files,
    packet_len,
    reduce,
    run_all,
    run_all_h16,
    run_all_h32,
    scheduled_elems,
    segment_count,
    segment_len,
    select_rounds,
    shuffle_h16,
)
