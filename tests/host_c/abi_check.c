/* Pure C99 consumer of include/ktanh.h: the header must compile as C, and the host-only entry
 * points must behave without a GPU.  Linked against libktanh.so by tests/test_boundary_host.py. */
#include <stdio.h>
#include <string.h>

#include "ktanh.h"

int main(void)
{
    const ktanh_lut_t *t1 = ktanh_default_lut();
    ktanh_lut_t fitted;
    ktanh_lut64_t fitted64;
    if (sizeof(ktanh_lut_t) != 96 || sizeof(ktanh_lut64_t) != 192) return 1;
    if (ktanh_lut_validate(t1) != KT_OK) return 2;
    if (ktanh_fit_lut(&fitted) != KT_OK || memcmp(&fitted, t1, sizeof fitted) != 0) return 3;
    if (ktanh_fit_lut64(&fitted64) != KT_OK || ktanh_lut64_validate(&fitted64) != KT_OK) return 4;
    if (ktanh_bf16(NULL, NULL, 0, NULL, NULL) != KT_OK) return 5;
    if (ktanh_bf16(NULL, NULL, 8, NULL, NULL) != KT_ERR_NULL) return 6;
    if (klstm_cell(NULL, NULL, NULL, NULL, 0, 1, 8, NULL, NULL) != KT_OK) return 7;
    fitted.r[3] = 9;
    if (ktanh_lut_validate(&fitted) != KT_ERR_LUT) return 8;
    printf("%s\n", ktanh_status_string(KT_OK));
    return 0;
}
