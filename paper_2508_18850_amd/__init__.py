"""Fused transformer decode block for AMD MI355X: thin binding over libcfdecode.so."""
from .binding import (CfConfig, CfError, DecodeBlock, algorithmic_bytes, decode_block_static, lib_path, load_library,  # noqa: F401
                      EXPORTED_SYMBOLS, TeamCollectives, TEAM_SUM, TEAM_MAX,
                      TEAM_ROUNDS, TEAM_TWO_KERNELS, TEAM_DIRECT, TEAM_TWO_HOPS, MlaBlock, MlaConfig, SplitHeadBlock,
                      FfnBlock, FfnConfig, FFN_SILU, FFN_GELU)
