/* A plain C99 client of the library: includes the header, links against libihip.so and calls the
 * entry points that need no GPU (version, workspace and slot arithmetic, argument checks and their
 * error text).  Built and run by tests/test_abi.py. */
#include <stdio.h>
#include <string.h>

#include "ihip.h"

int main(void)
{
    ihip_shape s;
    memset(&s, 0, sizeof s);
    s.B = 8; s.Hq = 32; s.Hkv = 8; s.d = 128; s.Tq = 1; s.b_q = 1;
    s.seq_lens = (const int32_t *)0x1000;           /* a device pointer the host never follows */
    s.max_seq_len = 1048576; s.n_sink = 128; s.n_stream = 1024;
    const int32_t chunks[4] = {256, 64, 16, 4}, keeps[4] = {256, 256, 512, 1024};
    printf("version %d\n", (int)ihip_version());
    printf("stage1_slots %d\n", (int)ihip_stage1_slots(&s, 256));
    printf("workspace %zu\n", ihip_workspace_bytes(IHIP_OP_DECODE_LAYER, &s, 4, chunks, keeps));
    ihip_tensor t = {0, 0, 0, 0};
    const int32_t rc = ihip_prune_stage(&s, t, t, 0, 0, 0, 256, 4092, 0, 0, 0);
    printf("null tensor rc %d: %s\n", (int)rc, ihip_last_error());
    s.d = 64;
    printf("d=64 rc %d\n", (int)ihip_stage1_slots(&s, 256));
    return 0;
}
