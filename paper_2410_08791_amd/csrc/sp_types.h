// Types shared by the host-side engine and the device code.
#pragma once
#include <stdint.h>

typedef uint16_t bf16_t;  // storage type for bfloat16 bit patterns
