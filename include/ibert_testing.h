/*
 * libibert -- hooks for tests and tuning runs.  Not part of the method and not needed by a user of the library:
 * nothing here changes a result.
 */
#ifndef IBERT_TESTING_H
#define IBERT_TESTING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Force tile configuration `config` (0 .. count-1) of the MFMA MatMul kernel for every later MatMul launch of this
 * process that takes the 16-byte aligned path; a negative value restores the built-in choice.  Returns the number of
 * configurations.  Process-wide and not thread-safe: for single-threaded tests that walk the kernel's instantiations
 * (Sec. 4.1's MatMuls are the same arithmetic under every tiling). */
int ibert_gemm_config_override(int32_t config);

/* Switch for A/B measurements: with `on` = 0 the MFMA MatMul gives each XCD a linear run of tiles instead of a near-square
 * block of the tile grid (the default, which fetches fewer operand bytes over the fabric).  Process-wide. */
void ibert_gemm_xcd_blocks(int32_t on);

/* While `device_word` (device uint32, owned by the caller) is non-NULL, every MFMA MatMul launch of this process has its
 * first workgroup store there which form of the epilogue it ran -- the choice depends on the per-channel shifts and
 * biases, which only the device sees.  NULL switches the record off.  Process-wide, not thread-safe. */
enum {
    IBERT_EPILOGUE_STAGED = 1,            /* through LDS, general 64-bit requantization, arithmetic GELU          */
    IBERT_EPILOGUE_DIRECT = 2,            /* register-direct (all shifts in [33, 62], |bias| < 2^30)              */
    IBERT_EPILOGUE_DIRECT_GELU_TABLE = 3, /* register-direct, GELU read from the workgroup's table in LDS         */
    IBERT_EPILOGUE_EDGE = 4               /* a tile on the edge of the output, or unaligned output rows           */
};
void ibert_gemm_epilogue_record(uint32_t* device_word);

#ifdef __cplusplus
}
#endif
#endif /* IBERT_TESTING_H */
