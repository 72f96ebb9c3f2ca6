// Return codes shared by the host-side sources (mirrors the enum in the public header).
#pragma once
#include "../../include/dla.h"
