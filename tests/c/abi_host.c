/* The boundary used from plain C (C99, no HIP headers): host packers, geometry, error codes.
 * Built and run by tests/test_host_lib.py; prints "ok" and returns 0 when every check holds. */
#include <stdio.h>
#include <string.h>

#include "tl.h"

int main(void)
{
    /* Sec. 3.1: code = w + 1, element 16 i + j in bits [2j+1 : 2j] of word i; a short row is padded with w = 0 */
    const int8_t w[1][20] = {{-1, 0, 1, 1, 0, -1, 1, 0, 0, 0, 1, -1, -1, 1, 0, 1, 1, -1, 0, 1}};
    uint32_t p2[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    int8_t back[1][20];
    uint32_t want0 = 0, want1 = 0;
    int j;
    for (j = 0; j < 16; ++j) want0 |= (uint32_t)(w[0][j] + 1) << (2 * j);
    for (j = 16; j < 32; ++j) want1 |= (uint32_t)((j < 20 ? w[0][j] : 0) + 1) << (2 * (j - 16));
    if (tl_row_stride_bytes(TL_FMT_2BIT, 20) != 8) return 1;
    if (tl_pack_2bit(&w[0][0], 1, 20, p2) != TL_OK) return 2;
    if (p2[0] != want0 || p2[1] != want1) return 3;
    if (tl_unpack(TL_FMT_2BIT, p2, 1, 20, &back[0][0]) != TL_OK) return 4;
    if (memcmp(back, w, sizeof w) != 0) return 5;
    /* Sec. 3.2 in its plain base-3 form: five weights per byte, sum (w_i + 1) 3^i */
    {
        uint8_t p3[16];
        memset(p3, 0xEE, sizeof p3);
        if (tl_row_stride_bytes(TL_FMT_1P6BIT, 20) != 16) return 6;
        if (tl_pack_1p6bit(&w[0][0], 1, 20, p3) != TL_OK) return 7;
        if (p3[0] != 0 + 1 * 3 + 2 * 9 + 2 * 27 + 1 * 81) return 8;
        if (tl_unpack(TL_FMT_1P6BIT, p3, 1, 20, &back[0][0]) != TL_OK) return 9;
        if (memcmp(back, w, sizeof w) != 0) return 10;
    }
    /* argument checks happen before anything touches a GPU */
    if (tl_pack_2bit(NULL, 1, 20, p2) != TL_ERR_NULL) return 11;
    if (tl_pack_2bit(&w[0][0], 0, 20, p2) != TL_ERR_SHAPE) return 12;
    if (tl_ternary_gemm(NULL, NULL, 0, NULL, 1, 1, 16, NULL) != TL_ERR_NULL) return 13;
    if (tl_status_str(TL_ERR_ALIGN) == NULL) return 14;
    printf("ok\n");
    return 0;
}
