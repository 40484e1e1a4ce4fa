/* Entry point of the sanitizer run of the C ABI's argument checks (tests/c_client). */
#include <stdio.h>
int duhl_c_client_argument_checks(void);
int main(void)
{
    const int rc = duhl_c_client_argument_checks();
    if (rc != 0) {
        fprintf(stderr, "argument check number %d failed\n", rc);
        return 1;
    }
    puts("C ABI argument checks under sanitizers: ok");
    return 0;
}
